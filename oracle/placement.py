"""Communication volume of a placement of data and computation blocks, written out from the definitions.
Test infrastructure (plain Python / numpy, nothing shared with the library).

Definitions followed:
  * Sec. 4.1: a computation block C_k = (Q_i, KV_j) consumes the data blocks Q_i and KV_j and contributes to O_i.
    Q, KV and O blocks of the same tokens live on the same device.  Total volume of a configuration:
        sum_k ( sum_{d in I_k} Size(d) [Dev(d) != Dev(C_k)] + sum_{o in O_k} Size(o) [Dev(o) != Dev(C_k)] ).
  * Sec. 4.2: hypergraph with one hyperedge per data block d, joining d to every computation block that consumes it
    or contributes to it, weight s_e = Size(d); connectivity metric  sum_e s_e (lambda_e - 1)  with lambda_e the
    number of devices the hyperedge's vertices span: each remote device moves the block once.
Here a table row is one computation block for all heads (the head dimension is not split), so Size(.) is the block's
token count times the bytes one token holds in that tensor (all heads).
"""
import numpy as np


def comm_volume(blk_len, table, blk_dev, comp_dev, n_devices, q_bytes, kv_bytes, o_bytes):
    """blk_len [n_blocks] tokens per block; table [n,3] (q_blk, kv_blk, kind; kind 3 = SKIP rows are not
    computation blocks); blk_dev [n_blocks], comp_dev [n] device ids.
    Returns dict(pairwise=Sec. 4.1 sum, connectivity=Sec. 4.2 metric, hyperedges=count of hyperedges with at
    least one computation block, send=[n_devices], recv=[n_devices] under the connectivity model)."""
    pairwise = 0
    q_users, kv_users, o_makers = {}, {}, {}
    for k, (qb, kb, kind) in enumerate(np.asarray(table).reshape(-1, 3).tolist()):
        if kind == 3:
            continue
        d = int(comp_dev[k])
        if blk_dev[qb] != d:
            pairwise += int(blk_len[qb]) * q_bytes       # fetch Q_i
            pairwise += int(blk_len[qb]) * o_bytes       # send the contribution to O_i
        if blk_dev[kb] != d:
            pairwise += int(blk_len[kb]) * kv_bytes      # fetch KV_j
        q_users.setdefault(qb, set()).add(d)
        kv_users.setdefault(kb, set()).add(d)
        o_makers.setdefault(qb, set()).add(d)
    conn = 0
    send = [0] * n_devices
    recv = [0] * n_devices
    edges = 0
    for users, per_token, outward in ((q_users, q_bytes, True), (kv_users, kv_bytes, True), (o_makers, o_bytes, False)):
        for b, devs in users.items():
            edges += 1
            owner = int(blk_dev[b])
            span = set(devs) | {owner}
            size = int(blk_len[b]) * per_token
            conn += size * (len(span) - 1)
            for d in span - {owner}:
                if outward:          # the owner sends the input block to d
                    send[owner] += size
                    recv[d] += size
                else:                # d sends its partial output to the owner
                    send[d] += size
                    recv[owner] += size
    return dict(pairwise=pairwise, connectivity=conn, hyperedges=edges, send=send, recv=recv)
