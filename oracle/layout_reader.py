"""Independent reader of the packed layouts (test infrastructure).

Written from the normative layout text in include/spqr.h, not from the
library's packer: it turns a packed byte buffer back into the logical arrays so
that the host packer can be checked on the CPU by a round trip.
"""
import numpy as np


def _pairs_from_dwords(dw, bits, npairs):
    """dw: uint32 [T, D] per-tile dwords -> (lo, hi) uint8 arrays [T, npairs]."""
    T = dw.shape[0]
    lo = np.zeros((T, npairs), dtype=np.uint8)
    hi = np.zeros((T, npairs), dtype=np.uint8)
    mask = (1 << bits) - 1
    for q in range(npairs):
        if bits == 4:
            d, off = q // 4, 4 * (q % 4)
            lo[:, q] = (dw[:, d] >> off) & mask
            hi[:, q] = (dw[:, d] >> (off + 16)) & mask
        else:
            t, e = q // 16, q % 16
            if e < 15:
                d, off = 3 * t + e // 5, 3 * (e % 5)
                lo[:, q] = (dw[:, d] >> off) & mask
                hi[:, q] = (dw[:, d] >> (off + 16)) & mask
            else:
                for i in range(3):
                    lo[:, q] |= (((dw[:, 3 * t + i] >> 15) & 1) << i).astype(np.uint8)
                    hi[:, q] |= (((dw[:, 3 * t + i] >> 31) & 1) << i).astype(np.uint8)
    return lo, hi


def read_packed(buf, m, n, w_bits, beta1, beta2, group_axis, layout_version=1):
    """Returns the logical arrays held by a packed uint8 buffer:
    layout 1: Q, s_q, z_q, s_s, z_s, s_z, z_z; layout 2: the same without s_z, z_z;
    layout 3: Q, s16, z16."""
    buf = np.ascontiguousarray(buf, dtype=np.uint8)
    tr_, tc_ = (beta2, beta1) if group_axis == 0 else (beta1, beta2)
    ntr, ntc = m // tr_, n // tc_
    kw = tr_ * tc_ * w_bits // 128
    nc = 3 * beta2 // 16                      # dwords of 3-bit statistic codes
    sd = {1: nc + 2, 2: nc + 1, 3: beta2}[layout_version]
    swf, sr = sd // 4, sd % 4
    tile_bytes = 16 * kw + 4 * sd
    assert buf.size == ntr * ntc * tile_bytes
    Q = np.zeros((m, n), dtype=np.uint8)
    gshape = (m, n // beta1) if group_axis == 0 else (m // beta1, n)
    s_q = np.zeros(gshape, dtype=np.uint16)   # 3-bit codes, or binary16 patterns for layout 3
    z_q = np.zeros(gshape, dtype=np.uint16)
    st2 = {k: np.zeros((ntr, ntc), dtype=np.uint16) for k in ("s_s", "z_s", "s_z", "z_z")}
    ppr = tc_ // 2
    for tr in range(ntr):
        for t0 in range(0, ntc, 64):
            L = min(64, ntc - t0)
            base = (tr * ntc + t0) * tile_bytes
            u32 = buf[base: base + L * tile_bytes].view(np.uint32)
            code = u32[: kw * L * 4].reshape(kw, L, 4).transpose(1, 0, 2).reshape(L, kw * 4)
            off = kw * L * 4
            full = u32[off: off + swf * L * 4].reshape(swf, L, 4).transpose(1, 0, 2).reshape(L, swf * 4)
            off += swf * L * 4
            rem = u32[off: off + sr * L].reshape(sr, L).T
            stat = np.concatenate([full, rem], axis=1)
            lo, hi = _pairs_from_dwords(code, w_bits, tr_ * ppr)
            tile = np.empty((L, tr_, tc_), dtype=np.uint8)
            tile[:, :, 0::2] = lo.reshape(L, tr_, ppr)
            tile[:, :, 1::2] = hi.reshape(L, tr_, ppr)
            Q[tr * tr_:(tr + 1) * tr_, t0 * tc_:(t0 + L) * tc_] = \
                tile.transpose(1, 0, 2).reshape(tr_, L * tc_)
            if layout_version == 3:  # dword g of the tile: s | z << 16
                sq, zq = stat & 0xFFFF, stat >> 16
            else:
                slo, shi = _pairs_from_dwords(stat, 3, beta2)
                seq = np.empty((L, 2 * beta2), dtype=np.uint8)
                seq[:, 0::2] = slo
                seq[:, 1::2] = shi
                sq, zq = seq[:, :beta2], seq[:, beta2:]
            if group_axis == 0:      # groups are the tile's rows: group grid [m, n/beta1]
                s_q[tr * tr_:(tr + 1) * tr_, t0:t0 + L] = sq.T
                z_q[tr * tr_:(tr + 1) * tr_, t0:t0 + L] = zq.T
            else:                    # groups are the tile's columns: group grid [m/beta1, n]
                s_q[tr, t0 * tc_:(t0 + L) * tc_] = sq.reshape(-1)
                z_q[tr, t0 * tc_:(t0 + L) * tc_] = zq.reshape(-1)
            if layout_version != 3:
                st2["s_s"][tr, t0:t0 + L] = stat[:, nc] & 0xFFFF
                st2["z_s"][tr, t0:t0 + L] = stat[:, nc] >> 16
            if layout_version == 1:
                st2["s_z"][tr, t0:t0 + L] = stat[:, nc + 1] & 0xFFFF
                st2["z_z"][tr, t0:t0 + L] = stat[:, nc + 1] >> 16
    if layout_version == 3:
        return dict(Q=Q, s16=s_q.view(np.float16), z16=z_q.view(np.float16))
    out = dict(Q=Q, s_q=s_q.astype(np.uint8), z_q=z_q.astype(np.uint8))
    keep = ("s_s", "z_s", "s_z", "z_z") if layout_version == 1 else ("s_s", "z_s")
    out.update({k: st2[k].view(np.float16) for k in keep})
    return out
