"""fp64 reference for spectral key editing and the causal attention that reads it.

TEST INFRASTRUCTURE: imported only by tests, the smoke check and the CPU-baseline
leg of the benchmark.  Shares no code, tables or helpers with the HIP kernels.

Every function takes and returns numpy float64 arrays (masks are integer arrays).
Shapes follow the key-editing hook of the paper's Algorithms 1 and 2:
keys are K[B, T, H, d] (batch, token, KV head, head dim) and the highlight mask
is m[B, T], shared by all heads.  Queries are Q[B, T, Hq, d] with Hq = G * H;
query head hq reads KV head hq // G (contiguous groups: a reading, the paper
does not state the grouping).

What is written out here, in the order the paper states it:

* Eq. 2            P = U_{:, :k} U_{:, :k}^T                      -> projector
* Sec. 3.3         P_dynamic = sum_m alpha_m U_m U_m^T            -> blended_projector
* Sec. 2 / Alg. 2  k' = k + g * P k on highlighted tokens only    -> edit_keys
* Eq. 2 + Eq. 4    k' = k + (g+ P+ k + g- P- k) / 2, P- from the trailing singular vectors
                                                                  -> edit_keys_eq4 (and eq4_as_low_rank:
                                                                     the same edit as a scaled key plus a
                                                                     signed low-rank update, fed to edit_keys)
* Sec. 2           Attn(i, j) = q_i . k_j / sqrt(d_k), causal softmax, weighted sum of V
                                                                  -> causal_attention
* Sec. 3.1         Omega = h^T h+- / n, SVD, smallest k with leading-singular-value mass >= gamma
                                                                  -> learn_projection
* Sec. 3.4         D_h = mean_i || h+_i - h-_i ||_2               -> head_relevance_distance
* generation step  the same attention for one new query per prompt over a cache of (edited) keys
                                                                  -> decode_attention
* query projection  Q[b,t,hq,:] = W_q[hq] x[b,t,:] (the linear map whose output the routing reads, Sec. 3.3)
                                                                  -> project_queries
* Eq. 6            alpha_m = sum_k (q.u_m^(k)) sigma_m^(k) / max_m |.|   -> route_eq6
* benchmark's routing rule  w = softmax_m(tau * cos(mean prompt query, prototype_m))
                                                                  -> route_softmax_cos

Pins (tests/test_oracle_*.py): closed form of Appendix C, score-side form of
Eq. 5, query-side form (Sec. 2), library scaled-dot-product attention,
brute-force scalar loops on tiny shapes, and for Eq. 4 the agreement of its two
independent forms plus its special cases (g- = 0, k- = d, hand-worked 2-d case).
No function here is unpinned.
"""
import numpy as np

_F = np.float64


def projector(U):
    """Eq. 2: orthogonal projector onto the span of the orthonormal columns of U[d, r]."""
    U = np.asarray(U, dtype=_F)
    return U @ U.T


def blended_projector(U_bank, alpha):
    """Sec. 3.3: P_dynamic = sum_m alpha_m * U_m U_m^T for one (layer, KV head).

    U_bank[M, d, r] holds the retained columns of every expert, alpha[M] the
    routing coefficients.  SEKA is the case M = 1, alpha = 1 (Appendix D).
    """
    U_bank = np.asarray(U_bank, dtype=_F)
    alpha = np.asarray(alpha, dtype=_F)
    d = U_bank.shape[1]
    P = np.zeros((d, d), dtype=_F)
    for m in range(U_bank.shape[0]):
        P += alpha[m] * projector(U_bank[m])
    return P


def edit_keys(K, U, gain, mask, w=None, key_scale=None):
    """Hook of Algorithms 1/2: K[b,t,h,:] = a_h * K[b,t,h,:] + g_h * P_{b,h} K[b,t,h,:] where m[b,t] != 0.

    K[B,T,H,d]; U[H,M,d,r]; gain[H] (0 = head not selected, Sec. 3.4);
    mask[B,T]; w[B,H,M] routing coefficients or None for all-ones (SEKA);
    key_scale[H] = a_h or None for 1 (a_h != 1 only arises from Eq. 4 with g- != 0, see eq4_as_low_rank).
    Returns a new array; rows that are not highlighted are copied untouched.
    """
    K = np.asarray(K, dtype=_F)
    U = np.asarray(U, dtype=_F)
    B, T, H, d = K.shape
    M = U.shape[1]
    K_out = K.copy()
    for b in range(B):
        hl = np.flatnonzero(np.asarray(mask[b]) != 0)
        if hl.size == 0:
            continue
        for h in range(H):
            g = float(gain[h])
            if g == 0.0:
                continue
            alpha = np.ones(M, dtype=_F) if w is None else np.asarray(w[b, h], dtype=_F)
            P = blended_projector(U[h], alpha)
            k = K[b, hl, h, :]                      # [n, d], one key per row
            delta = g * (k @ P.T)                   # row form of g * P k
            a = 1.0 if key_scale is None else float(key_scale[h])
            K_out[b, hl, h, :] = a * k + delta
    return K_out


def edit_keys_eq4(K, U_pos, U_neg, k_pos, k_neg, g_pos, g_neg, mask):
    """Eq. 2 and Eq. 4 written out: k' = k + (g+ P+ k + g- P- k) / 2 on highlighted tokens, with
    P+ = U+[:, :k+] U+[:, :k+]^T (leading singular vectors) and P- = U-[:, k-:] U-[:, k-:]^T (trailing ones).

    K[B,T,H,d]; U_pos, U_neg [H,d,d] full sets of left singular vectors (orthogonal matrices);
    k_pos, k_neg [H] integers; g_pos, g_neg scalars or [H]; mask[B,T].
    """
    K = np.asarray(K, dtype=_F)
    B, T, H, d = K.shape
    gp = np.broadcast_to(np.asarray(g_pos, dtype=_F), (H,))
    gn = np.broadcast_to(np.asarray(g_neg, dtype=_F), (H,))
    K_out = K.copy()
    for h in range(H):
        Up = np.asarray(U_pos[h], dtype=_F)[:, :int(k_pos[h])]
        Un = np.asarray(U_neg[h], dtype=_F)[:, int(k_neg[h]):]
        P_pos = Up @ Up.T
        P_neg = Un @ Un.T
        for b in range(B):
            hl = np.flatnonzero(np.asarray(mask[b]) != 0)
            k = K[b, hl, h, :]
            K_out[b, hl, h, :] = k + (gp[h] * (k @ P_pos.T) + gn[h] * (k @ P_neg.T)) / 2.0
    return K_out


def eq4_as_low_rank(U_pos, U_neg, k_pos, k_neg, g_pos, g_neg, B):
    """Eq. 4 in the form the hook takes.  Because U- is orthogonal, its trailing columns project onto the
    complement of its leading ones: P- = I - U-[:, :k-] U-[:, :k-]^T, so
        k' = (1 + g-/2) k + (g+/2) U+[:, :k+] U+[:, :k+]^T k - (g-/2) U-[:, :k-] U-[:, :k-]^T k,
    i.e. two "experts" per head (leading k+ columns of U+, leading k- columns of U-, zero-padded to one
    width r = max(k+, k-) rounded up to a multiple of 8), gain 1, coefficients (g+/2, -g-/2), key scale 1 + g-/2.
    Returns U[H,2,d,r], gain[H], w[B,H,2], key_scale[H].
    """
    H, d, _ = np.asarray(U_pos).shape
    gp = np.broadcast_to(np.asarray(g_pos, dtype=_F), (H,))
    gn = np.broadcast_to(np.asarray(g_neg, dtype=_F), (H,))
    r = int(max(max(int(x) for x in k_pos), max(int(x) for x in k_neg), 1))
    r = (r + 7) // 8 * 8
    U = np.zeros((H, 2, d, r), dtype=_F)
    for h in range(H):
        U[h, 0, :, :int(k_pos[h])] = np.asarray(U_pos[h], dtype=_F)[:, :int(k_pos[h])]
        U[h, 1, :, :int(k_neg[h])] = np.asarray(U_neg[h], dtype=_F)[:, :int(k_neg[h])]
    w = np.zeros((B, H, 2), dtype=_F)
    w[:, :, 0] = gp / 2.0
    w[:, :, 1] = -gn / 2.0
    return U, np.ones(H, dtype=_F), w, 1.0 + gn / 2.0


def causal_attention(Q, K, V, scale=None):
    """Sec. 2: scores q_i.k_j / sqrt(d_k) for j <= i, softmax over j, weighted sum of V.

    Materialises the full T x T score matrix per (batch, query head).
    Returns O[B,T,Hq,d] and LSE[B,Hq,T] (log of the softmax denominator,
    including the subtracted row maximum).
    """
    Q = np.asarray(Q, dtype=_F)
    K = np.asarray(K, dtype=_F)
    V = np.asarray(V, dtype=_F)
    B, T, Hq, d = Q.shape
    H = K.shape[2]
    G = Hq // H
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    O = np.empty_like(Q)
    LSE = np.empty((B, Hq, T), dtype=_F)
    visible = np.tril(np.ones((T, T), dtype=bool))
    for b in range(B):
        for hq in range(Hq):
            h = hq // G
            A = scale * (Q[b, :, hq, :] @ K[b, :, h, :].T)       # [T, T]
            A = np.where(visible, A, -np.inf)
            row_max = A.max(axis=1, keepdims=True)
            E = np.exp(A - row_max)
            denom = E.sum(axis=1, keepdims=True)
            O[b, :, hq, :] = (E / denom) @ V[b, :, h, :]
            LSE[b, hq, :] = (row_max + np.log(denom))[:, 0]
    return O, LSE


def steered_attention(Q, K, V, U, gain, mask, w=None, scale=None, key_scale=None):
    """Edited keys first (materialised), then ordinary causal attention on them."""
    K_edit = edit_keys(K, U, gain, mask, w, key_scale)
    return causal_attention(Q, K_edit, V, scale)


def attention_rows(Q, K, V, rows, scale=None):
    """The same attention for a list of (b, hq, i) output rows, one at a time.

    K is whatever the queries should see (already edited if steering is on).
    Each row only needs keys and values 0..i, so this is how outputs are
    checked at sizes where the full score matrix is too large for the host.
    Returns O_rows[n, d] and LSE_rows[n].
    """
    B, T, Hq, d = Q.shape
    H = K.shape[2]
    G = Hq // H
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    out = np.empty((len(rows), d), dtype=_F)
    lse = np.empty(len(rows), dtype=_F)
    for n, (b, hq, i) in enumerate(rows):
        h = hq // G
        q = np.asarray(Q[b, i, hq, :], dtype=_F)
        k = np.asarray(K[b, : i + 1, h, :], dtype=_F)
        v = np.asarray(V[b, : i + 1, h, :], dtype=_F)
        a = scale * (k @ q)
        a_max = a.max()
        e = np.exp(a - a_max)
        s = e.sum()
        out[n] = (e / s) @ v
        lse[n] = a_max + np.log(s)
    return out, lse


def decode_attention(q, K, V, lens=None, scale=None):
    """Generation step after the prompt (the edited keys persist in the KV cache, Algorithm 1's hook ran at
    prefill): one new query per (prompt, head) attends to the first lens[b] cached keys, its own included.

    q[B,Hq,d]; K, V [B,Tmax,H,d] caches (K already edited where the prompt was highlighted);
    lens[B] number of valid cached tokens per prompt, or None for Tmax.
    Returns O[B,Hq,d] and LSE[B,Hq].
    """
    q = np.asarray(q, dtype=_F)
    B, Hq, d = q.shape
    H = K.shape[2]
    G = Hq // H
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    O = np.empty((B, Hq, d), dtype=_F)
    LSE = np.empty((B, Hq), dtype=_F)
    for b in range(B):
        n = K.shape[1] if lens is None else int(lens[b])
        for hq in range(Hq):
            h = hq // G
            k = np.asarray(K[b, :n, h, :], dtype=_F)
            v = np.asarray(V[b, :n, h, :], dtype=_F)
            a = scale * (k @ q[b, hq])
            a_max = a.max()
            e = np.exp(a - a_max)
            O[b, hq] = (e / e.sum()) @ v
            LSE[b, hq] = a_max + np.log(e.sum())
    return O, LSE


def learn_projection(h_neutral, h_signal, gamma):
    """Offline spectral learning for one layer (Sec. 3.1): per KV head, the cross-covariance
    Omega = h^T h_signal / n of token key embeddings, its SVD Omega = U S V^T, and the smallest k whose
    leading singular values hold at least a fraction gamma of their sum.

    h_neutral, h_signal [n, H, d].  Returns U[H,d,d] (columns = left singular vectors, singular values
    descending), S[H,d], k[H] (1 <= k <= d).  Eq. 2 then takes U[:, :k] (positive side) or U[:, k:] (negative).
    """
    hn = np.asarray(h_neutral, dtype=_F)
    hs = np.asarray(h_signal, dtype=_F)
    n, H, d = hn.shape
    U = np.empty((H, d, d), dtype=_F)
    S = np.empty((H, d), dtype=_F)
    k = np.empty(H, dtype=np.int64)
    for h in range(H):
        omega = hn[:, h, :].T @ hs[:, h, :] / n
        u, sv, _ = np.linalg.svd(omega)
        U[h], S[h] = u, sv
        frac = np.cumsum(sv) / sv.sum()
        k[h] = int(np.searchsorted(frac, gamma - 1e-15) + 1)
        k[h] = min(max(k[h], 1), d)
    return U, S, k


def head_relevance_distance(h_pos, h_neg):
    """Sec. 3.4: D_h = mean over tokens of || h+_i - h-_i ||_2, per KV head.  h_pos, h_neg [n, H, d]."""
    diff = np.asarray(h_pos, dtype=_F) - np.asarray(h_neg, dtype=_F)
    return np.sqrt((diff * diff).sum(axis=-1)).mean(axis=0)


def mean_group_query(Q, H, t0, t1):
    """Mean of the queries of tokens [t0, t1) over the G query heads of each KV head.

    Q[B,T,Hq,d] -> q_bar[B,H,d].  [t0, t1) = [T-1, T) is the paper's last-token
    query (Sec. 3.3); [0, T) is the benchmark's mean prompt query.
    """
    Q = np.asarray(Q, dtype=_F)
    B, T, Hq, d = Q.shape
    G = Hq // H
    q_bar = np.empty((B, H, d), dtype=_F)
    for b in range(B):
        for h in range(H):
            q_bar[b, h] = Q[b, t0:t1, h * G:(h + 1) * G, :].reshape(-1, d).mean(axis=0)
    return q_bar


def project_queries(X, Wq, Hq):
    """Q[b, t, hq, d] = sum_e X[b, t, e] Wq[hq * D + d, e]: the layer's query projection, one weight row per
    output feature (paper Sec. 3.3 routes on these queries)."""
    X = np.asarray(X, dtype=np.float64)
    Wq = np.asarray(Wq, dtype=np.float64)
    B, T, E = X.shape
    N = Wq.shape[0]
    assert Wq.shape[1] == E and N % Hq == 0
    Q = np.zeros((B, T, N))
    for n in range(N):                      # one output feature at a time: a dot product per token
        Q[:, :, n] = X @ Wq[n]
    return Q.reshape(B, T, Hq, N // Hq)


def route_softmax_cos(Q, proto, t0, t1, tau):
    """Benchmark routing rule: w = softmax_m(tau * cos(q_bar, prototype_m)).

    proto[H,M,d].  A zero-length q_bar or prototype gives cos = 0 for that
    expert (so all-zero queries give uniform weights).  Returns w[B,H,M].
    """
    proto = np.asarray(proto, dtype=_F)
    H, M, d = proto.shape
    q_bar = mean_group_query(Q, H, t0, t1)
    B = q_bar.shape[0]
    w = np.empty((B, H, M), dtype=_F)
    for b in range(B):
        for h in range(H):
            cos = np.zeros(M, dtype=_F)
            qn = np.sqrt(q_bar[b, h] @ q_bar[b, h])
            for m in range(M):
                pn = np.sqrt(proto[h, m] @ proto[h, m])
                if qn * pn >= 1e-30:
                    cos[m] = (q_bar[b, h] @ proto[h, m]) / (qn * pn)
            z = tau * cos
            e = np.exp(z - z.max())
            w[b, h] = e / e.sum()
    return w


def route_eq6(Q, U_top, sigma, t0, t1):
    """Eq. 6: alpha_m = sum_{k<=K} (q.u_m^(k)) sigma_m^(k) / max_m' |sum_k ...|.

    U_top[H,M,d,K] are the top-K left singular vectors of every expert,
    sigma[H,M,K] their singular values.  q is the query of tokens [t0, t1)
    averaged over the query heads of the group (the paper uses the last
    token, [T-1, T)).  If every alignment is below 1e-30 in magnitude the
    coefficients are 0 (no steering).  Returns alpha[B,H,M].
    """
    U_top = np.asarray(U_top, dtype=_F)
    sigma = np.asarray(sigma, dtype=_F)
    H, M, d, Ktop = U_top.shape
    q_bar = mean_group_query(Q, H, t0, t1)
    B = q_bar.shape[0]
    alpha = np.zeros((B, H, M), dtype=_F)
    for b in range(B):
        for h in range(H):
            a = np.zeros(M, dtype=_F)
            for m in range(M):
                for k in range(Ktop):
                    a[m] += (q_bar[b, h] @ U_top[h, m, :, k]) * sigma[h, m, k]
            biggest = np.abs(a).max()
            if biggest >= 1e-30:
                alpha[b, h] = a / biggest
    return alpha
