"""A hand-worked two-step, three-layer run of the expansion stage (paper, "Dynamic Expansion
Stage": Eq. 1, Eq. 2, Algorithm 1, the depth-pruning buffers), shared by the oracle pin and the
native parity test.  Every expected number below was worked out on paper from the definitions;
none comes from running either implementation.

Grid L = 4, M = 3, one sample per batch (Eq. 1's average is then the prefix sum), prompt n0 = 2,
C1 = 0.24, C2 = 0.48, buffers of R = 2 values.

Tables (row r is the context (r+1)*L; Eq. 2 divides the draft row by the target's first entry):
  row 0: S_D = 1 2 3 4, S_T[.][1] = 1  ->  c = 1    2   3    4
  row 1: S_D = 1 2 3 4, S_T[.][1] = 2  ->  c = 0.5  1   1.5  2
  row 2: S_D = 1 2 3 4, S_T[.][1] = 4  ->  c = 0.25 0.5 0.75 1

Step 1.
  layer 1: context 2 -> row 0.  v = .8 .4 .3 .1, u = .8 1.2 1.5 1.6.  Chords into 4: from 2 it is
           .4/2 = .2 < C1, so 4 is invalid; into 3: .35, .3; into 2: .4.  n_1 = 3, u = 1.5, c = 3.
           alpha_1 = 1: 1 * 1.5/3 = .5 >= C2, go on.
  layer 2: context 2 + 3 = 5 -> row 1 (with the context stuck at 2 it would be row 0, where the
           chord 2 -> 3 is .125/1 < C1 and only 2 nodes would be kept).  v = .5 .25 .125 .1,
           u = .5 .75 .875 .975.  Chords: 1->2 .5, 2->3 .25, 1->3 .375, 3->4 .2 < C1.  n_2 = 3,
           u = .875, c = 1.5.  phi_1 = .875/1.5 = 7/12 goes into A_1 = {1, 7/12}.
           alpha_2 = 1: .875/1.5 = .58333 >= C2, go on.  (Had phi_1 been put into A_2, alpha_2 would
           be 19/24 and 19/24 * 7/12 = .4618 < C2: the step would stop at two layers.)
  layer 3: context 8 -> row 2.  v = .6 .2 .04 .02, u = .6 .8 .84 .86.  Chords: 1->2 .8,
           2->3 .04/.25 = .16 < C1, 3->4 .08 < C1.  n_3 = 2, u = .8, c = .5.
           phi_2 = .8/.875 = 32/35 goes into A_2 = {1, 32/35}.  Last layer offered: no test.
  kept = 3 3 2; alpha_1 = 19/24, alpha_2 = 67/70, alpha_3 = 1.

Step 2 (same buffers).
  layer 1: row 0.  v = .9 .6 .5 .1, u = .9 1.5 2.0 2.1.  Chord 3->4 is .1 < C1; the others are
           >= .5.  n_1 = 3, u = 2, c = 3.  alpha_1 * 2/3 = 19/36 = .5278 >= C2, go on.
  layer 2: context 5 -> row 1.  v = .3 .19 .01 .01, u = .3 .49 .5 .51.  Chords: 1->2 .38,
           2->3 .02 < C1, 3->4 .02 < C1, 2->4 .02 < C1.  n_2 = 2, u = .49, c = 1.
           phi_1 = .49/2 = .245 goes into A_1, which drops its oldest value: A_1 = {7/12, .245}.
           alpha_2 * .49/1 = 67/70 * .49 = .469 < C2: stop (with a fresh buffer .49 >= C2 would go on).
  kept = 3 2; alpha_1 = (7/12 + .245)/2, alpha_2 = 67/70.
"""
L, M, N0, C1, C2, R = 4, 3, 2, 0.24, 0.48, 2
S_D = [[1.0, 2.0, 3.0, 4.0]] * 3
S_T = [[1.0, 1.5, 2.0, 2.5], [2.0, 2.5, 3.0, 3.5], [4.0, 4.5, 5.0, 5.5]]
STEP1 = [[[0.8, 0.4, 0.3, 0.1]], [[0.5, 0.25, 0.125, 0.1]], [[0.6, 0.2, 0.04, 0.02]]]
STEP2 = [[[0.9, 0.6, 0.5, 0.1]], [[0.3, 0.19, 0.01, 0.01]], [[0.6, 0.2, 0.04, 0.02]]]
KEPT1, KEPT2 = [3, 3, 2], [3, 2]
ALPHA_AFTER_1 = {1: 19.0 / 24.0, 2: 67.0 / 70.0, 3: 1.0}
ALPHA_AFTER_2 = {1: (7.0 / 12.0 + 0.245) / 2.0, 2: 67.0 / 70.0, 3: 1.0}
BUFFERS_AFTER_1 = {1: [1.0, 7.0 / 12.0], 2: [1.0, 32.0 / 35.0]}
BUFFERS_AFTER_2 = {1: [7.0 / 12.0, 0.245], 2: [1.0, 32.0 / 35.0]}
