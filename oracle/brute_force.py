"""Scalar brute force of the LM head for tiny shapes (test infrastructure, not product).

Pure-Python loops over Python floats (IEEE double): no array library, no shared helpers with
the vectorised oracle.  Forward is Eq. 1 written out element by element; backward is the
per-(b,v) update of Alg. 3 with the derivative of log(1+ReLU(x)) taken as 1/(1+x).
Same readings as the oracle: the mask excludes positions, lowest index wins ties, a row without
valid tokens gives 0 / index 0 / no gradient, the gate is strict.
"""
import math


def forward(H, W, bias, mask):
    B, S, D, V = len(H), len(H[0]), len(H[0][0]), len(W)
    Y = [[0.0] * V for _ in range(B)]
    I = [[0] * V for _ in range(B)]
    X = [[-math.inf] * V for _ in range(B)]
    for b in range(B):
        for v in range(V):
            best_act = 0.0     # Eq. 1: masked positions contribute exactly 0 to the max
            have_any = False
            for s in range(S):
                logit = bias[v]
                for d in range(D):
                    logit += H[b][s][d] * W[v][d]
                act = math.log1p(logit if logit > 0.0 else 0.0) * (1.0 if mask[b][s] else 0.0)
                if act > best_act:
                    best_act = act
                if mask[b][s] and (not have_any or logit > X[b][v]):
                    X[b][v] = logit
                    I[b][v] = s
                    have_any = True
            Y[b][v] = best_act
    return Y, I, X


def backward(H, W, bias, mask, dY):
    B, S, D, V = len(H), len(H[0]), len(H[0][0]), len(W)
    _, I, X = forward(H, W, bias, mask)
    dH = [[[0.0] * D for _ in range(S)] for _ in range(B)]
    dW = [[0.0] * D for _ in range(V)]
    db = [0.0] * V
    for b in range(B):
        for v in range(V):
            x = X[b][v]
            if not (x > 0.0):
                continue
            g = dY[b][v] / (1.0 + x)
            s = I[b][v]
            db[v] += g
            for d in range(D):
                dW[v][d] += g * H[b][s][d]
                dH[b][s][d] += g * W[v][d]
    return dH, dW, db
