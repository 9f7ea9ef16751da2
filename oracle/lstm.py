"""CPU oracle for the ONNX LSTM operator (test infrastructure only): the operator's equations
evaluated step by step in double precision with numpy.  Nothing here is used by the GPU
library, and nothing here uses it.  (The paper names LSTM among the operators its compiler
supports, Section 4.1, and leaves the arithmetic to the ONNX standard.)

Definition (default activations, no peepholes, layout 0).  X [seq, batch, input];
W [dirs, 4H, input], R [dirs, 4H, H] with the gate blocks in the order i, o, f, c along the 4H
axis; B [dirs, 8H] = the four input biases followed by the four recurrent biases in the same
order; initial_h, initial_c [dirs, batch, H] (zeros when absent).  For each direction and time
step t (time runs backwards for the reverse direction):

    i = sigmoid(x_t Wi' + h Ri' + Wbi + Rbi)        f = sigmoid(x_t Wf' + h Rf' + Wbf + Rbf)
    g = tanh   (x_t Wc' + h Rc' + Wbc + Rbc)        o = sigmoid(x_t Wo' + h Ro' + Wbo + Rbo)
    c = f * c + i * g                               h = o * tanh(c)

Y [seq, dirs, batch, H] collects h of every step at its time index, Y_h and Y_c [dirs, batch, H]
are the last h and c of each direction.
"""
import numpy as np


def _sigmoid(v):
    return 1.0 / (1.0 + np.exp(-v))


def lstm(X, W, R, B=None, initial_h=None, initial_c=None, direction="forward"):
    X = np.asarray(X, dtype=np.float32).astype(np.float64)
    W = np.asarray(W, dtype=np.float32).astype(np.float64)
    R = np.asarray(R, dtype=np.float32).astype(np.float64)
    seq, batch, _ = X.shape
    dirs = {"forward": 1, "reverse": 1, "bidirectional": 2}[direction]
    H = R.shape[2]
    assert W.shape[0] == dirs and R.shape[0] == dirs and W.shape[1] == 4 * H and R.shape[1] == 4 * H
    Bv = np.zeros((dirs, 8 * H)) if B is None else np.asarray(B, dtype=np.float32).astype(np.float64)
    h0 = np.zeros((dirs, batch, H)) if initial_h is None else np.asarray(initial_h, dtype=np.float32).astype(np.float64)
    c0 = np.zeros((dirs, batch, H)) if initial_c is None else np.asarray(initial_c, dtype=np.float32).astype(np.float64)
    Y = np.zeros((seq, dirs, batch, H))
    Yh = np.zeros((dirs, batch, H))
    Yc = np.zeros((dirs, batch, H))
    for d in range(dirs):
        backwards = direction == "reverse" or d == 1
        Wi, Wo, Wf, Wc = (W[d, k * H:(k + 1) * H] for k in range(4))
        Ri, Ro, Rf, Rc = (R[d, k * H:(k + 1) * H] for k in range(4))
        bi, bo, bf, bc = (Bv[d, k * H:(k + 1) * H] + Bv[d, (4 + k) * H:(5 + k) * H] for k in range(4))
        h, c = h0[d].copy(), c0[d].copy()
        for step in range(seq):
            t = seq - 1 - step if backwards else step
            x = X[t]
            i = _sigmoid(x @ Wi.T + h @ Ri.T + bi)
            f = _sigmoid(x @ Wf.T + h @ Rf.T + bf)
            g = np.tanh(x @ Wc.T + h @ Rc.T + bc)
            o = _sigmoid(x @ Wo.T + h @ Ro.T + bo)
            c = f * c + i * g
            h = o * np.tanh(c)
            Y[t, d] = h
        Yh[d], Yc[d] = h, c
    return Y, Yh, Yc
