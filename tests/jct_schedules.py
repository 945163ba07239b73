"""Hand-worked schedules of the job-completion-time model (bulk-synchronous training under
stragglers; Section II Eq. 1, Section VI-A steps 1-5, Section VII-A.2/3).

Every expected value below is a literal worked out by hand from the rules as the header of the
library states them (and Section VI-A gives them); none was produced by running the oracle or
the library.  All quantities are small integers or dyadic fractions, so every comparison is
exact in double precision.  The same cases check the oracle (tests/test_oracle_pins.py) and the
library (tests/test_host_logic.py).

Rules used:  T_i = t0_i + B_i / v_i + delay_i;  an iteration takes max_i T_i + t_server;
decisions at the first iteration end at or after each multiple of decide_every;  window means
over the iterations that ended within the last L seconds;  slow trigger (Section VI-A step 3):
max_i mean T_i >= lambda * mean over workers;  v_i = mean of B_i / T_i over the window;  Eq. 3
split: the integer split that minimises max_i B_i / v_i;  kill (Section VI-A step 4): the slowest
worker over L_per when >= lambda * mean, absent for restart_cost seconds, back without its
persistent delay, no batch-size decision at that decision;  equal split whenever the set of
present workers changes;  BACKUP_WORKERS (Section VII-A.3): the b slowest of an iteration are
disregarded, their samples do not count.
"""
BSP, ADJUST_BS, BACKUP_WORKERS, ANTDT_ND = 0, 1, 2, 3

SCHEDULES = []


def _case(name, cfg, **expected):
    SCHEDULES.append((name, cfg, expected))


# A. ADJUST_BS by the slow-worker rule of Section VI-A step 3.  Two workers, 1 sample/s each,
#    worker 1 carries a persistent delay of 18 s.
#    it 1: sizes [6, 6]; T = [6, 6 + 18 = 24]; ends at t = 24 (< 40: no decision)
#    it 2: the same; ends at t = 48 >= 40 -> decision.  Window (60 s) holds both iterations:
#          mean T = [6, 24], their mean 15; 24 >= 1.5 * 15 = 22.5 -> ADJUST_BS.
#          v = [6/6, 6/24] = [1, 1/4].  Eq. 3 for B = 12: (10, 2) costs max(10, 8) = 10;
#          (9, 3) costs 12; (11, 1) costs 11 -> sizes [10, 2].
#    it 3: T = [10, 2 + 18 = 20]; ends at t = 68.  36 samples done: the job ends.
_case("adjust_bs_slow_worker",
      dict(n=2, B=12, N=36, t0=[0.0, 0.0], v=[1.0, 1.0], persistent_delay=[0.0, 18.0], policy=ADJUST_BS,
           decide_every=40.0, L_trans=60.0, L_per=60.0, lam=1.5),
      jct=68.0, iterations=3, processed=36, adjust_actions=1, kills=0, max_bpt=24.0, sum_bpt=68.0,
      final_sizes=[10, 2])

# B. KILL_RESTART of a persistent straggler (Section VI-A step 4) with a server term of 1 s.
#    Three workers, 1 sample/s, worker 2 delayed by 20 s; restart takes 30 s.
#    it 1-2: sizes [4, 4, 4]; T = [4, 4, 24]; each iteration 24 + 1 = 25 s -> t = 25, 50.
#    t = 50 >= 50 -> decision: mean T over L_per = [4, 4, 24], their mean 32/3; 24 >= 1.5 * 32/3 = 16
#          -> worker 2 is killed, absent until 50 + 30 = 80; no batch-size decision now.
#    it 3-7: workers {0, 1}, equal split [6, 6]; 6 + 1 = 7 s each -> t = 57, 64, 71, 78, 85
#          (iteration 7 starts at 78 < 80: worker 2 is still away).
#    it 8-10: started at 85 >= 80: worker 2 is back, without its delay; equal split [4, 4, 4];
#          4 + 1 = 5 s each -> t = 90, 95, 100.
#    t = 100 >= 100 -> decision: means over the last 100 s: workers 0, 1: (4+4 + 5*6 + 3*4)/10 = 5,
#          worker 2 (history restarted): 4; their mean 14/3; 5 < 1.5 * 14/3 = 7: nobody is killed;
#          5 < 7 and 4 * 1.5 = 6 > 14/3: no ADJUST_BS.  120 samples done: the job ends.
#    sum of batch times = 2*24 + 5*6 + 3*4 = 90; plus ten server terms = 100.
_case("kill_restart_persistent_straggler",
      dict(n=3, B=12, N=120, t0=[0.0] * 3, v=[1.0] * 3, t_server=1.0, persistent_delay=[0.0, 0.0, 20.0],
           policy=ANTDT_ND, decide_every=50.0, L_trans=100.0, L_per=100.0, lam=1.5, restart_cost=30.0),
      jct=100.0, iterations=10, processed=120, adjust_actions=0, kills=1, max_bpt=24.0, sum_bpt=90.0,
      final_sizes=[4, 4, 4])

# C. The same cluster under plain BSP and under BACKUP_WORKERS with b = 1 (Section VII-A.3).
#    BSP: ten iterations of 24 + 1 s.  Backup workers: worker 2 is dropped every iteration, which
#    then takes 4 + 1 s and completes 8 samples: 15 iterations for 120 samples.
_case("bsp_paced_by_the_straggler",
      dict(n=3, B=12, N=120, t0=[0.0] * 3, v=[1.0] * 3, t_server=1.0, persistent_delay=[0.0, 0.0, 20.0],
           policy=BSP),
      jct=250.0, iterations=10, processed=120, adjust_actions=0, kills=0, max_bpt=24.0, sum_bpt=240.0,
      final_sizes=[4, 4, 4])
_case("backup_workers_drop_the_straggler",
      dict(n=3, B=12, N=120, t0=[0.0] * 3, v=[1.0] * 3, t_server=1.0, persistent_delay=[0.0, 0.0, 20.0],
           policy=BACKUP_WORKERS, backup_b=1),
      jct=75.0, iterations=15, processed=120, adjust_actions=0, kills=0, max_bpt=4.0, sum_bpt=60.0,
      final_sizes=[4, 4, 4])

# D. Burst bookkeeping of Section VII-A.2 with every (window, worker) pair disturbed (prob = 1,
#    so the pseudo-random choice plays no part): bursts are the first 10 s of every 20 s; a
#    disturbed iteration is 2 * 1.5 = 3 s longer; whether an iteration is disturbed is decided
#    when it starts.  Two workers, B = 8, 1 sample/s: an iteration takes 4 s, or 7 s in a burst.
#    starts 0 (burst) -> 7; 7 (burst) -> 14; 14 -> 18; 18 -> 22; 22 (2 s into the second
#    period: burst) -> 29; 29 (9 s: burst) -> 36; 36 -> 40.  Seven iterations, 56 samples.
_case("bursts_delay_the_iterations_that_start_inside_them",
      dict(n=2, B=8, N=56, t0=[0.0, 0.0], v=[1.0, 1.0], period=20.0, duration=10.0, prob=1.0,
           sleep_duration=2.0, intensity=1.5, seed=5, policy=BSP),
      jct=40.0, iterations=7, processed=56, adjust_actions=0, kills=0, max_bpt=7.0, sum_bpt=40.0,
      final_sizes=[4, 4])

# E. The window decides whether a second ADJUST_BS comes.  True speeds [1, 1/4] samples/s, no
#    delays, lambda = 1.2, decisions every 30 s.
#    it 1: sizes [10, 10]; T = [10, 40]; t = 40 >= 30 -> decision: mean 25; 40 >= 30 -> ADJUST_BS,
#          v = [1, 1/4]; Eq. 3 for B = 20: (16, 4) costs 16 on both sides, any other split more.
#    it 2-3: T = [16, 16]; t = 56, 72.  t = 72 >= 60 -> decision.
#      window 40 s: iterations that ended after t = 32, i.e. at 40, 56, 72: mean T =
#          [(10+16+16)/3, (40+16+16)/3] = [14, 24], their mean 19; 24 >= 1.2 * 19 = 22.8 ->
#          ADJUST_BS again (v = [1, 1/4] in all three iterations: the split stays [16, 4]).
#      window 20 s: iterations that ended after t = 52, i.e. at 56, 72: mean T = [16, 16]:
#          no straggler (16 < 19.2) and no fast worker (16 * 1.2 > 16): no action.
_E = dict(n=2, B=20, N=60, t0=[0.0, 0.0], v=[1.0, 0.25], policy=ADJUST_BS, decide_every=30.0, L_per=100.0, lam=1.2)
_case("window_still_holds_the_unbalanced_iteration", dict(_E, L_trans=40.0),
      jct=72.0, iterations=3, processed=60, adjust_actions=2, kills=0, max_bpt=40.0, sum_bpt=72.0,
      final_sizes=[16, 4])
_case("window_holds_balanced_iterations_only", dict(_E, L_trans=20.0),
      jct=72.0, iterations=3, processed=60, adjust_actions=1, kills=0, max_bpt=40.0, sum_bpt=72.0,
      final_sizes=[16, 4])

# F. The added trigger (a reading that goes beyond Section VI-A: a worker lambda times FASTER
#    than the mean also starts ADJUST_BS, so that a worker whose disturbance has ended gets its
#    share back).  Two workers, worker 1 delayed by 6 s: T = [6, 12], mean 9; the slow rule does
#    not fire (12 < 13.5), the fast rule does (6 * 1.5 = 9 <= 9).
#    it 1-2: t = 12, 24 >= 20 -> decision -> v = [1, 1/2]; Eq. 3 for B = 12: (8, 4) costs 8 on both
#          sides.  it 3: T = [8, 4 + 6 = 10]; t = 34.
_case("fast_worker_trigger_reading",
      dict(n=2, B=12, N=36, t0=[0.0, 0.0], v=[1.0, 1.0], persistent_delay=[0.0, 6.0], policy=ADJUST_BS,
           decide_every=20.0, L_trans=60.0, L_per=60.0, lam=1.5),
      jct=34.0, iterations=3, processed=36, adjust_actions=1, kills=0, max_bpt=12.0, sum_bpt=34.0,
      final_sizes=[8, 4])

# G. The slow-worker rule of Section VI-A step 3 alone (the added fast-worker trigger does not
#    fire here).  Three workers, 1 sample/s, worker 2 delayed by 5 s: T = [4, 4, 9], mean 17/3;
#    9 >= 1.5 * 17/3 = 8.5 (slow rule), 4 * 1.5 = 6 > 17/3 (no fast worker).
#    it 1-2: t = 9, 18 >= 15 -> decision -> v = [1, 1, 4/9].  Eq. 3 for B = 12: (5, 5, 2) costs
#          max(5, 5, 2 * 9/4 = 4.5) = 5; every other split costs more ((5, 4, 3): 6.75; (6, 4, 2): 6).
#    it 3: T = [5, 5, 2 + 5 = 7]; t = 25.
_case("slow_rule_without_the_fast_trigger",
      dict(n=3, B=12, N=36, t0=[0.0] * 3, v=[1.0] * 3, persistent_delay=[0.0, 0.0, 5.0], policy=ADJUST_BS,
           decide_every=15.0, L_trans=60.0, L_per=60.0, lam=1.5),
      jct=25.0, iterations=3, processed=36, adjust_actions=1, kills=0, max_bpt=9.0, sum_bpt=25.0,
      final_sizes=[5, 5, 2])
