"""CPU oracle of the locality-preserving block rearrange (App. "Rearrange for Locality Preserving", Alg. 3).

Test infrastructure: only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline may use it.  It shares
no code with the HIP path.  The function is the algorithm's three steps as printed there -- reshape into
(N_t, B_t, N_h, B_h, N_w, B_w, .), permute to (N_t, N_h, N_w, B_t, B_h, B_w, .), flatten to (N_b, B, .) --
followed by what the cache layout adds and the paper leaves to the implementation: the feature dimension
d = heads x d_h is split and the heads moved to the front, because every head has its own cache."""
import numpy as np


def blockify(X, Bt, Bh, Bw):
    """X [T][Hs][Ws][H][d] (any dtype) -> [H][N_b][Bt*Bh*Bw][d]."""
    T, Hs, Ws, H, d = X.shape
    assert T % Bt == 0 and Hs % Bh == 0 and Ws % Bw == 0, "Alg. 3 assumes exact division"
    Nt, Nh, Nw = T // Bt, Hs // Bh, Ws // Bw
    x = X.reshape(Nt, Bt, Nh, Bh, Nw, Bw, H, d)            # group into blocks
    x = x.transpose(0, 2, 4, 1, 3, 5, 6, 7)                # block-contiguous layout
    x = x.reshape(Nt * Nh * Nw, Bt * Bh * Bw, H, d)        # flatten to block-major
    return np.ascontiguousarray(x.transpose(2, 0, 1, 3))   # one cache per head


def unblockify(Xb, T, Hs, Ws, Bt, Bh, Bw):
    """[H][N_b][Bt*Bh*Bw][d] -> [T][Hs][Ws][H][d]: the steps of blockify undone in reverse order."""
    H, Nb, B, d = Xb.shape
    Nt, Nh, Nw = T // Bt, Hs // Bh, Ws // Bw
    x = Xb.transpose(1, 2, 0, 3).reshape(Nt, Nh, Nw, Bt, Bh, Bw, H, d)
    x = x.transpose(0, 3, 1, 4, 2, 5, 6, 7)
    return np.ascontiguousarray(x.reshape(T, Hs, Ws, H, d))
