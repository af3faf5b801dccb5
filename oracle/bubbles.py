"""Bubble model: where one GPU's share of a distributed training step idles, and for how long.

The paper observes bubbles (Sec. 2.1 "Idle GPU Computing Resources": communication waits in DP and MP,
pipeline bubbles in PP) but gives no formula; on one GPU they are modelled as waits of a length derived from
the bytes a collective would move at a fixed bandwidth (DP, TP) or from the 1F1B schedule (PP).  All times are
integer nanoseconds, bytes * 1e9 // bandwidth (floor).

A bubble list is a list of (site, ns): `site` names the position in the step's kernel sequence after which the
training stream idles.
"""


def collective_ns(n_bytes, bw_bytes_per_s):
    return (int(n_bytes) * 1_000_000_000) // int(bw_bytes_per_s)


def dp_bubbles(n_params, bytes_per_grad, bw_bytes_per_s, ring_factor_num=1, ring_factor_den=1,
               exposed_num=1, exposed_den=1):
    """Data parallel: one exposed gradient all-reduce after backward, before the optimizer.

    Literal reading of the configuration: time = gradient bytes / bandwidth.  ring_factor (2(N-1)/N for a
    ring) and the exposed fraction (1 - overlap with backward) default to 1.
    """
    g = n_params * bytes_per_grad
    ns = collective_ns(g * ring_factor_num * exposed_num, bw_bytes_per_s * ring_factor_den * exposed_den)
    return [("after_backward", ns)]


def tp_bubbles(n_layers, tokens, d_model, bytes_per_act, bw_bytes_per_s):
    """Tensor parallel (Megatron-style): an activation all-reduce after the two row-parallel GEMMs of each
    layer in forward (attention out-projection, MLP down-projection) and after the two column-parallel
    dgrads in backward (QKV, MLP up-projection): 4 per layer per step, each tokens*d_model*bytes long."""
    ns = collective_ns(tokens * d_model * bytes_per_act, bw_bytes_per_s)
    out = []
    for l in range(n_layers):
        out.append((f"fwd{l}.attn_out", ns))
        out.append((f"fwd{l}.mlp_down", ns))
    for l in reversed(range(n_layers)):
        out.append((f"bwd{l}.mlp_up_dgrad", ns))
        out.append((f"bwd{l}.qkv_dgrad", ns))
    return out


def pp_1f1b_ops(stage, n_stages, n_micro):
    """Order in which a 1F1B stage runs its forward (F,k) and backward (B,k) passes: p-1-s warm-up forwards,
    then alternating one forward / one backward, then the remaining backwards."""
    w = min(n_stages - 1 - stage, n_micro)
    ops = [("F", k) for k in range(w)]
    f, b = w, 0
    while f < n_micro:
        ops.append(("F", f)); f += 1
        ops.append(("B", b)); b += 1
    while b < n_micro:
        ops.append(("B", b)); b += 1
    return ops


def pp_1f1b_bubbles(stage, n_stages, n_micro, t_f_ns, t_b_ns):
    """Idle intervals of one 1F1B stage with uniform forward time t_f and backward time t_b per micro-batch
    (n_micro >= n_stages).  Returns [(site, ns)], site = ("before", op) for a gap in front of that op or
    ("end", None) for the wait until the slowest stage finishes.  Zero-length gaps are omitted.
    Total = (p-1)(t_f+t_b) for every stage."""
    assert n_micro >= n_stages
    s, p = stage, n_stages
    w = p - 1 - s
    out = []
    if s > 0:
        out.append((("before", ("F", 0)), s * t_f_ns))
    if w > 0:
        out.append((("before", ("B", 0)), w * t_b_ns))
        for k in range(n_micro - w, n_micro):
            out.append((("before", ("B", k)), t_f_ns))
    if s > 0:
        out.append((("end", None), s * t_b_ns))
    return out


def dp_gradient_buckets(group_bytes, cap_bytes):
    """Data parallel with bucketed gradient exchange (a reading beyond the configuration's single exposed
    all-reduce; Sec. 2.1 only says that communication leaves the GPU idle).

    `group_bytes[i]` = gradient bytes that become final together, listed in the order in which backward
    finalizes them.  Groups are appended to the open bucket; the bucket is closed as soon as it holds at least
    `cap_bytes` (so a group larger than the cap closes the bucket it joins), and whatever is open at the end
    forms the last bucket.  Returns a list of buckets, each a list of group indices.
    """
    assert cap_bytes > 0
    buckets, cur, held = [], [], 0
    for i, b in enumerate(group_bytes):
        cur.append(i)
        held += int(b)
        if held >= cap_bytes:
            buckets.append(cur)
            cur, held = [], 0
    if cur:
        buckets.append(cur)
    return buckets


def dp_overlapped_wait(ready_ns, dur_ns, end_ns):
    """Exposed wait of a bucketed all-reduce that runs beside backward.

    Bucket k can be sent once its gradients are final (`ready_ns[k]`) and the bucket before it has been sent (one
    exchange at a time, in bucket order); sending it takes `dur_ns[k]`.  Backward ends at `end_ns`, and the
    optimizer has to wait until the last bucket has arrived: the wait is what is left of the exchange then, zero
    if it is already over.  Integer nanoseconds throughout.
    """
    assert len(ready_ns) == len(dur_ns)
    finish = 0
    for r, d in zip(ready_ns, dur_ns):
        start = max(int(r), finish)
        finish = start + int(d)
    return max(0, finish - int(end_ns))
