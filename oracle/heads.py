"""Loss head and embedding optimiser of the training step, NumPy.  TEST INFRASTRUCTURE ONLY (see the package docstring).

The paper's training loop (Section 2: the forward pass ends in a loss, its gradients update the model parameters and,
for learnable base representations, the lookup table) names neither the node-classification loss nor the optimiser.
Readings taken here:
  - node classification: softmax cross-entropy of the encoder's output row against the node's class label;
  - learnable base representations: Adagrad per element (accumulate the squared gradient, divide the step by the
    root of the accumulator), as an alternative to the plain SGD of embedding_sgd.
"""
import numpy as np


def softmax_xent(logits: np.ndarray, labels: np.ndarray, grad_scale: float = 1.0):
    """loss[i] = logsumexp(logits[i]) - logits[i, labels[i]];  grad[i] = grad_scale * (softmax(logits[i]) - onehot),
    the gradient of grad_scale * sum(loss) with respect to the logits.  fp64."""
    z = np.asarray(logits, dtype=np.float64)
    labels = np.asarray(labels, dtype=np.int64)
    m = z.max(axis=1, keepdims=True)
    e = np.exp(z - m)
    s = e.sum(axis=1, keepdims=True)
    lse = (m + np.log(s))[:, 0]
    loss = lse - z[np.arange(len(labels)), labels]
    grad = e / s
    grad[np.arange(len(labels)), labels] -= 1.0
    return loss, grad * float(grad_scale)


def embedding_adagrad(table: np.ndarray, state: np.ndarray, node_ids: np.ndarray, d_h0: np.ndarray, lr: float,
                      eps: float):
    """Adagrad on the rows of the lookup table that the batch touched, in fp32 with every operation rounded on its own:
        state[v] += g * g;   table[v] -= lr * g / (sqrt(state[v]) + eps)      for v = node_ids[r], g = d_h0[r].
    node_ids holds every node once.  Returns updated copies (table, state)."""
    t = np.array(table, dtype=np.float32, copy=True)
    s = np.array(state, dtype=np.float32, copy=True)
    g = np.asarray(d_h0, dtype=np.float32)
    acc = s[node_ids] + g * g
    s[node_ids] = acc
    step = (np.float32(lr) * g) / (np.sqrt(acc) + np.float32(eps))
    t[node_ids] = t[node_ids] - step
    return t, s


def mean_xent_grad(logits: np.ndarray, labels: np.ndarray) -> np.ndarray:
    """d(mean over the rows of the softmax cross-entropy)/d(logits), stored as fp32: the upstream gradient dL/dH^k
    that the tests, the smoke check and the benchmark's CPU leg hand to the backward pass of both sides."""
    return softmax_xent(logits, labels, 1.0 / len(labels))[1].astype(np.float32)
