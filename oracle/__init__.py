"""CPU oracle for the PPO / BC / symmetry / RND hot path and its recurrent variant (fp64, numpy).

TEST INFRASTRUCTURE ONLY.  This package is a plain, slow, obviously-correct
statement of what the GPU library computes.  It is imported by the tests, by
the smoke check and by the benchmark's CPU-baseline leg, and by nothing else:
the product path never calls it and shares no code, tables or helpers with it.

Everything is computed in float64 from the caller's (float32) inputs.  Library
primitives used as steps: numpy matmul, numpy stable argsort.  There is no
blocking, fusion or reordering beyond what each cited definition states.

Pin status (what independent fact each function is checked against lives in
tests/test_oracle_*.py):
  rng.mix64 / permutation / act_noise ... pinned (big-int reimplementation,
                                          bijection, moments)
  gae.gae ............................... pinned (closed forms, O(T^2) brute force)
  gae.normalize_advantages .............. pinned (mean 0, unbiased std 1)
  gaussian.* ............................ pinned (scipy normal pdf, entropy closed form,
                                          Monte-Carlo KL)
  mlp.forward / backward ................ pinned (affine special case, finite differences)
  ppo.minibatch_loss_and_grads .......... pinned (ratio==1 case, clip cases,
                                          finite differences of the scalar loss)
  adam.clip_scale / adam.adam_step ...... pinned (hand-stepped scalar table)
  symmetry.* ............................ pinned (involution, equivariant net, identity map)
  bc.* .................................. pinned (zero loss, normal-equation gradient)
  rnd.* ................................. pinned (two-pass mean/var, zero error)
  gru.cell / sequence_forward ........... pinned (library GRU cell and GRU in fp64, closed forms,
                                          separately run episodes for the resets)
  gru.cell_backward / sequence_backward . pinned (finite differences, library autodiff, per-episode
                                          brute force)
  lstm.cell / sequence_forward / cell_backward / sequence_backward
                                          pinned (library LSTM cell and LSTM in fp64, closed forms,
                                          per-episode brute force, finite differences, library autodiff)
  recurrent.* with cell="lstm" .......... pinned (on-policy identities, finite differences of both losses)
  recurrent.act / minibatch_loss_and_grads / ppo_update
                                          pinned (act == sequence re-run, on-policy identities, finite
                                          differences of the scalar loss, column-wise minibatches)
  recurrent.bc_collect_step / bc_minibatch_loss_and_grad / bc_update
                                          pinned (zero loss on the student's own roll-out, finite
                                          differences, memory-free special case == bc.bc_loss_and_grad)
"""
