"""CPU oracle for the polybasic speculative-decoding verify path.

TEST INFRASTRUCTURE ONLY.  Plain, slow, fp64 implementations of what the GPU
path computes, written from the paper's definitions; nothing in the product
package imports this, and this imports nothing from the product package.

  accept.py / accept.c   speculative-sampling acceptance (VERIFY of Algorithm 1)
  forward.py             decoder-only transformer forward pass, M_i(x_{<=t})
  chain.py               Algorithm 1 generalised to an n-level chain
  theory.py              Eq. (2), Lemma 3.1, Theorem 3.2, Theorem 3.3 closed forms
"""
