"""Row-sampled and any-size checks of the training step (TEST INFRASTRUCTURE ONLY).

For partitions too large for the whole-step oracle, each function here evaluates the paper's
definition (Eq. 1-2 and the chain rule on them) for a handful of rows, columns or relations,
in float64 NumPy, from given layer inputs.  A dense matmul is the only library step.  Every
function is pinned against the whole-step C oracle on a small graph (tests/test_oracle_sampled.py).
"""
from __future__ import annotations

import numpy as np


class EdgeView:
    """Per-edge arrays of a partition in its sorted order: destination, relation, 1/c_{i,r}."""

    def __init__(self, part):
        lens = np.diff(part["seg_ptr"])
        seg = np.repeat(np.arange(part["n_seg"]), lens)
        self.src = part["col_src"]
        self.dst = part["seg_dst"][seg]
        self.rel = part["seg_rel"][seg]
        self.invc = (1.0 / lens.astype(np.float64))[seg]
        self.n_vert = part["n_vert"]

    def into(self, rows):
        """Edge indices whose destination is in `rows`."""
        mask = np.zeros(self.n_vert, bool); mask[np.asarray(rows)] = True
        return np.nonzero(mask[self.dst])[0]

    def out_of(self, rows):
        mask = np.zeros(self.n_vert, bool); mask[np.asarray(rows)] = True
        return np.nonzero(mask[self.src])[0]


def project_rows(H_rows, V):
    """P[j][b][:] = h_j V_b for the given rows (Eq. 2 applied to h_j).  H_rows [n, d_in]."""
    return np.einsum("nk,bko->nbo", np.asarray(H_rows, np.float64), np.asarray(V, np.float64))


def transposed_rows(ev: EdgeView, rows, a, G):
    """dP[j][b][:] = sum over edges j -> i under r of a_rb (1/c_{i,r}) G_i, for sources `rows`.
    G is the full [N, d] gradient with respect to the pre-activations (any float dtype)."""
    a = np.asarray(a, np.float64)
    rows = np.asarray(rows)
    B, d = a.shape[1], G.shape[1]
    out = np.zeros((len(rows), B, d))
    e = ev.out_of(rows)
    slot = {int(j): k for k, j in enumerate(rows)}
    for idx in e:
        g = np.asarray(G[ev.dst[idx]], np.float64)
        out[slot[int(ev.src[idx])]] += (a[ev.rel[idx]] * ev.invc[idx])[:, None] * g[None, :]
    return out


def input_grad_rows(dP_rows, G_rows, V, W0):
    """dH_j = sum_b dP[j][b][:] V_b^T + G_j W_0^T  (chain rule on h_j V_b and h_j W_0)."""
    V = np.asarray(V, np.float64); W0 = np.asarray(W0, np.float64)
    return (np.einsum("nbo,bko->nk", np.asarray(dP_rows, np.float64), V)
            + np.asarray(G_rows, np.float64) @ W0.T)


def self_weight_grad(H_in, G, chunk=1 << 18):
    """dW_0 = H^T G over all vertices, accumulated in float64 chunk by chunk."""
    d_in, d_out = H_in.shape[1], G.shape[1]
    out = np.zeros((d_in, d_out))
    for s in range(0, H_in.shape[0], chunk):
        g = np.asarray(G[s:s + chunk], np.float64)
        nz = np.nonzero(np.abs(g).max(axis=1) > 0)[0]
        if len(nz):
            out += np.asarray(H_in[s:s + chunk][nz], np.float64).T @ g[nz]
    return out


def basis_weight_grad_column(H_in, dP_col, chunk=1 << 20):
    """dV_b[:, c] = H^T dP[:, b, c]: one column of one basis gradient, from that column of dP."""
    out = np.zeros(H_in.shape[1])
    for s in range(0, H_in.shape[0], chunk):
        out += np.asarray(H_in[s:s + chunk], np.float64).T @ np.asarray(dP_col[s:s + chunk], np.float64)
    return out


def coeff_grad_relations(ev: EdgeView, rels, P_of, G, B):
    """da[r][b] = sum over edges j -> i under r of (1/c_{i,r}) <P[j][b][:], G_i>, for the listed
    relations.  P_of(src_ids) returns the projected rows [n, B, d] of those sources."""
    out = {}
    for r in rels:
        e = np.nonzero(ev.rel == r)[0]
        acc = np.zeros(B)
        for s in range(0, len(e), 256):
            ee = e[s:s + 256]
            P = np.asarray(P_of(ev.src[ee]), np.float64)
            g = np.asarray(G[ev.dst[ee]], np.float64)
            acc += np.einsum("e,ebo,eo->b", ev.invc[ee], P, g)
        out[int(r)] = acc
    return out


def euler_quantity(pre, H_in, W0, G, chunk=1 << 18):
    """Q = sum_i <pre_i - h_i W_0, G_i>.  Because the aggregate is linear in the coefficients and in
    the bases, Q = sum_{r,b} a_rb da_rb = sum_b <dV_b, V_b>  at any size.  `pre` only has to be
    right where G is non-zero (so ReLU outputs serve as pre-activations there)."""
    q = 0.0
    W0 = np.asarray(W0, np.float64)
    for s in range(0, G.shape[0], chunk):
        g = np.asarray(G[s:s + chunk], np.float64)
        nz = np.nonzero(np.abs(g).max(axis=1) > 0)[0]
        if len(nz):
            agg = np.asarray(pre[s:s + chunk][nz], np.float64) - np.asarray(H_in[s:s + chunk][nz], np.float64) @ W0
            q += float(np.sum(agg * g[nz]))
    return q


# ---- the regrouped evaluation of Eq. 1-2 (run means z, per-basis sums y), sampled ----------------
def run_mean_rows(part, runs, H):
    """z_s = (1/c_s) sum_{j in run s} h_j for the listed runs."""
    out = np.zeros((len(runs), H.shape[1]))
    for k, s in enumerate(runs):
        src = part["col_src"][part["seg_ptr"][s]:part["seg_ptr"][s + 1]]
        out[k] = np.asarray(H[src], np.float64).sum(0) / len(src)
    return out


def basis_sum_rows(part, rows, a, Z_of):
    """y_{i,b} = sum over the runs (r, i) of destination i of a_rb z_{(r,i)}, for destinations `rows`.
    Z_of(run_ids) returns the stored run means of those runs [n, d]."""
    a = np.asarray(a, np.float64)
    order = np.argsort(part["seg_dst"], kind="stable")
    first = np.searchsorted(part["seg_dst"][order], rows, "left")
    last = np.searchsorted(part["seg_dst"][order], rows, "right")
    out = []
    for f, l in zip(first, last):
        runs = order[f:l]
        z = np.asarray(Z_of(runs), np.float64) if len(runs) else np.zeros((0, 1))
        out.append(np.einsum("sb,sk->bk", a[part["seg_rel"][runs]], z) if len(runs) else None)
    d = next((o.shape[1] for o in out if o is not None), 1)
    return np.stack([o if o is not None else np.zeros((a.shape[1], d)) for o in out])


def coeff_grad_relations_runs(part, rels, Z_of, V, G):
    """da[r][b] = sum over the runs s = (r, i) of relation r of <z_s V_b, G_i>  (the chain rule on
    y_{i,b} = sum_r a_rb z_{i,r}, pre_i = sum_b y_{i,b} V_b + ...), for the listed relations."""
    V = np.asarray(V, np.float64)
    out = {}
    for r in rels:
        runs = np.nonzero(part["seg_rel"] == r)[0]
        acc = np.zeros(V.shape[0])
        for s in range(0, len(runs), 512):
            rr = runs[s:s + 512]
            z = np.asarray(Z_of(rr), np.float64)
            g = np.asarray(G[part["seg_dst"][rr]], np.float64)
            acc += np.einsum("sk,bkc,sc->b", z, V, g)
        out[int(r)] = acc
    return out


def transposed_column(ev: EdgeView, a, b, G_col):
    """dP[:, b, col] for every source: sum over its out-edges of a_rb (1/c) G[dst][col], given column
    `col` of G as a vector over vertices."""
    a = np.asarray(a, np.float64)
    w = a[ev.rel, b] * ev.invc * np.asarray(G_col, np.float64)[ev.dst]
    return np.bincount(ev.src, weights=w, minlength=ev.n_vert)


def relation_weight(a, V, r):
    """W_r = sum_b a_rb V_b (Eq. 2)."""
    return np.einsum("b,bkc->kc", np.asarray(a, np.float64)[r], np.asarray(V, np.float64))


def relation_product_rows(part, runs, Z_of, a, V):
    """u_s = z_s W_{rel(s)} for the listed runs (z as Z_of returns it)."""
    z = np.asarray(Z_of(runs), np.float64)
    out = np.zeros((len(runs), np.shape(V)[2]))
    for k, s in enumerate(runs):
        out[k] = z[k] @ relation_weight(a, V, part["seg_rel"][s])
    return out


def relation_product_t_rows(part, runs, G, a, V):
    """dz_s = G_{dst(s)} W_{rel(s)}^T for the listed runs (chain rule on u_s = z_s W_r)."""
    out = np.zeros((len(runs), np.shape(V)[1]))
    for k, s in enumerate(runs):
        out[k] = np.asarray(G[part["seg_dst"][s]], np.float64) @ relation_weight(a, V, part["seg_rel"][s]).T
    return out


# ---- reductions over every vertex or edge, at any size ----------------------------------------------
def basis_weight_grad_projection(ev: EdgeView, a, H_in, G, x, y):
    """x^T dV_b y for every basis b, where dV_b = H^T dP_b and dP[j][b][:] = sum over edges j -> i under r
    of a_rb (1/c_{i,r}) G_i (chain rule on Eq. 1-2):
        x^T dV_b y = sum_e (h_{src(e)} . x) a_{rel(e), b} (1/c_e) (G_{dst(e)} . y)
    One pass over the edges whatever the sizes; checks every element of dV_b in one random direction."""
    a = np.asarray(a, np.float64)
    hx = np.asarray(H_in, np.float64) @ np.asarray(x, np.float64)        # [N]
    gy = np.asarray(G, np.float64) @ np.asarray(y, np.float64)           # [N]
    w = hx[ev.src] * ev.invc * gy[ev.dst]                                # one term per edge
    per_rel = np.bincount(ev.rel, weights=w, minlength=a.shape[0])       # sum over the edges of a relation
    return per_rel @ a                                                   # [B]


def coeff_grad_relation_edges(ev: EdgeView, r, H_in, G, V, chunk=1 << 18):
    """da[r][b] for every basis b of ONE relation, however many edges it has:
        da_rb = sum over edges j -> i under r of (1/c_{i,r}) <h_j V_b, G_i> = <C_r, V_b>,
        C_r = sum_e (1/c_e) h_{src(e)}^T G_{dst(e)}     (d_in x d_out, a dense product chunk by chunk)."""
    V = np.asarray(V, np.float64)
    live = np.zeros(ev.n_vert, bool)                 # edges into rows whose gradient is zero add nothing
    for s in range(0, ev.n_vert, 1 << 20):
        live[s:s + (1 << 20)] = np.abs(G[s:s + (1 << 20)]).max(axis=1) > 0
    e = np.nonzero((ev.rel == r) & live[ev.dst])[0]
    C = np.zeros(V.shape[1:])
    for s in range(0, len(e), chunk):
        ee = e[s:s + chunk]
        g = np.asarray(G[ev.dst[ee]], np.float64) * ev.invc[ee][:, None]
        C += np.asarray(H_in[ev.src[ee]], np.float64).T @ g
    return np.einsum("kc,bkc->b", C, V)
