"""Oracle: the versatile-workload policy as pure integer logic (test infrastructure only).

Follows Sec. 4.3 (roles, Eq. 1, policy boundary), the Record step of Alg. 2 (census,
boundary predicate, spare promotion), Alg. 6 (policy_adjustment), Alg. 7
(policy_advancement) and Alg. 8 (the adaptive strawman).  Notation is the paper's:
W_init, G_init, B = W_init * G_init, W_cur, G_cur, R_cur, C_cur, G_ext, eps (world epoch).

Readings taken where the paper leaves a choice (each is listed in the design notes):
  * roles after advancement go to survivors in ascending original index: majors, the
    minor, major-spares, minor-spares (agrees with the Sec. 4.3 example, where r29 of 31
    is the minor and r31 the minor-spare);
  * the boundary minors are the LAST n_bdry contributing survivors in ascending order;
  * spares stay masked at a boundary and are left out of C_cur and of the W that sizes
    G_ext, so that Eq. 1 can always be met exactly;
  * a vacated slot is filled by the lowest-index spare of the same role whose quota
    equals the lost quota (always the case between boundaries);
  * quotas ("targets") are totals for the iteration; the extension is sized from the
    quota deficit B - sum(target of contributing survivors), which at the synchronisation
    point (where the paper detects failures) equals B - C_cur.
"""

MAJOR, MINOR, MAJOR_SPARE, MINOR_SPARE, DEAD = 0, 1, 2, 3, 4
RESTORE_SKIP, RESTORE_BLOCKING, RESTORE_NONBLOCKING = 0, 1, 2


class NoSurvivor(Exception):
    """Every replica has failed; the guarantee needs one survivor (Sec. 4, Claim)."""


def smallest_G_cur(W_cur, B):
    """Alg. 7, choice of G_cur: count G up until W_cur * G >= B."""
    G = 1
    while W_cur * G < B:
        G += 1
    return G


def smallest_G_ext(C_cur, W_cur, B):
    """Alg. 6 boundary branch: count G_ext up from 1 until C_cur + W_cur * G_ext >= B."""
    G_ext = 1
    while C_cur + W_cur * G_ext < B:
        G_ext += 1
    return G_ext


def policy_advancement(W_cur, B):
    """Alg. 7: steady-state layout for W_cur survivors.

    Returns dict(G_cur, n_maj, n_min, R_cur, n_ms, n_mi).
    """
    G_cur = smallest_G_cur(W_cur, B)
    n_maj = B // G_cur
    R_cur = B - n_maj * G_cur
    n_min = 1 if R_cur > 0 else 0
    spare = W_cur - n_maj - n_min
    n_mi = 1 if (n_min == 1 and spare >= 2) else 0
    n_ms = spare - n_mi
    return dict(G_cur=G_cur, n_maj=n_maj, n_min=n_min, R_cur=R_cur, n_ms=n_ms, n_mi=n_mi)


def boundary_extension(C_cur, W_cur, B):
    """Alg. 6 boundary branch: (G_ext, n_bdry)."""
    G_ext = smallest_G_ext(C_cur, W_cur, B)
    n_bdry = W_cur * G_ext - (B - C_cur)
    return G_ext, n_bdry


class World:
    """Role, quota and epoch bookkeeping of one cross-replica group.

    static=True is the paper's StaticWorldPolicy; static=False is Alg. 8.
    """

    def __init__(self, W_init, G_init, static=True):
        assert W_init >= 1 and G_init >= 1
        self.W_init, self.G_init = W_init, G_init
        self.B = W_init * G_init
        self.static = static
        self.role = [MAJOR] * W_init
        self.G_cur, self.R_cur = G_init, 0
        self.eps = 0
        self.pending_advance = False
        self.begin_iteration()

    # ---- views -------------------------------------------------------------------
    def alive(self):
        return [r for r in range(self.W_init) if self.role[r] != DEAD]

    def contributors(self):
        """Survivors whose buffers enter the reduction: majors and minors (Alg. 2, Reduce)."""
        return [r for r in range(self.W_init) if self.role[r] in (MAJOR, MINOR)]

    def quota_of_role(self, role):
        if role in (MAJOR, MAJOR_SPARE):
            return self.G_cur
        if role in (MINOR, MINOR_SPARE):
            return self.R_cur
        return 0

    def role_counts(self):
        bm = self.is_boundary_minor
        n = lambda k: sum(1 for r in range(self.W_init) if self.role[r] == k and not bm[r])
        return dict(n_maj=n(MAJOR), n_min=n(MINOR), n_ms=n(MAJOR_SPARE), n_mi=n(MINOR_SPARE),
                    n_bm=sum(1 for r in self.alive() if bm[r]))

    # ---- iteration lifecycle -----------------------------------------------------
    def begin_iteration(self):
        """Alg. 1, start of the iteration: counters to zero, quotas from the roles (Sec. 4.3)."""
        W = self.W_init
        self.contributed = [0] * W
        self.target = [self.quota_of_role(self.role[r]) for r in range(W)]
        self.is_boundary_minor = [False] * W
        self.loop_bound = self.G_cur              # P(major)
        self.crossed_boundary = False
        self.restore_mode = RESTORE_SKIP

    def should_contribute(self, r):
        """Alg. 1, quota test: accumulate while the quota is not met."""
        return self.role[r] != DEAD and self.contributed[r] < self.target[r]

    def C_cur(self):
        return sum(self.contributed[r] for r in self.contributors())

    def committed_total(self):
        return self.C_cur()

    # ---- failure inside an iteration ---------------------------------------------
    def on_failure(self, failed):
        """Record (Alg. 2) + handle_work_failure (Alg. 4) + policy_adjustment (Alg. 6 / 8)."""
        failed = sorted(set(failed))
        assert failed, "on_failure needs a non-empty failure set"
        for r in failed:
            assert 0 <= r < self.W_init and self.role[r] != DEAD
        if len(failed) == len(self.alive()):
            raise NoSurvivor()
        lost = [(self.role[r], self.target[r]) for r in failed]
        for r in failed:                          # Repair: shrink to the survivors
            self.role[r] = DEAD
            self.is_boundary_minor[r] = False
        self.eps += 1

        G_ext = n_bdry = 0
        if not self.static:                       # Alg. 8: repair and continue
            at_boundary = False
            self.restore_mode = RESTORE_BLOCKING
        else:
            unfilled = 0
            for role, quota in lost:              # Record: promote or declare a boundary
                if role not in (MAJOR, MINOR):
                    continue                      # a lost spare vacates no slot
                want = MAJOR_SPARE if role == MAJOR else MINOR_SPARE
                cand = [s for s in self.alive() if self.role[s] == want and self.target[s] == quota]
                if cand:
                    self.role[cand[0]] = role
                else:
                    unfilled += 1
            at_boundary = unfilled > 0
            if not at_boundary:                   # Alg. 6, non-boundary branch
                self.restore_mode = RESTORE_BLOCKING
            else:                                 # Alg. 6, boundary branch
                con = self.contributors()
                W_c = len(con)
                if W_c == 0:                      # only spares left: they take over as majors
                    for s in self.alive():
                        self.role[s] = MAJOR if self.role[s] == MAJOR_SPARE else MINOR
                    con = self.contributors()
                    W_c = len(con)
                planned = sum(self.target[r] for r in con)
                G_ext, n_bdry = boundary_extension(planned, W_c, self.B)
                for k, r in enumerate(con):
                    if k >= W_c - n_bdry:
                        self.target[r] += G_ext - 1
                        self.is_boundary_minor[r] = True
                    else:
                        self.target[r] += G_ext
                for s in self.alive():            # spares keep shadowing a full major/minor
                    if self.role[s] in (MAJOR_SPARE, MINOR_SPARE):
                        self.target[s] += G_ext
                self.loop_bound += G_ext
                self.crossed_boundary = True
                self.restore_mode = RESTORE_NONBLOCKING
        return self.decision(at_boundary, G_ext, n_bdry)

    def decision(self, at_boundary=False, G_ext=0, n_bdry=0):
        d = dict(at_boundary=int(at_boundary), restore_mode=self.restore_mode, epoch=self.eps,
                 W_cur=len(self.alive()), C_cur=self.C_cur(), G_ext=G_ext, n_bdry=n_bdry,
                 G_cur=self.G_cur, R_cur=self.R_cur, loop_bound=self.loop_bound,
                 role=list(self.role), target=list(self.target),
                 contributed=list(self.contributed),
                 is_boundary_minor=[int(x) for x in self.is_boundary_minor])
        d.update(self.role_counts())
        return d

    # ---- commit ------------------------------------------------------------------
    def commit(self):
        """Alg. 1's commit step has run; start the next iteration's counters."""
        self.pending_advance = self.crossed_boundary
        self.begin_iteration()

    def advance(self):
        """Alg. 1 after the commit / Alg. 7: only after an iteration that crossed a boundary."""
        if self.pending_advance:
            lay = policy_advancement(len(self.alive()), self.B)
            self.G_cur, self.R_cur = lay["G_cur"], lay["R_cur"]
            seq = ([MAJOR] * lay["n_maj"] + [MINOR] * lay["n_min"] +
                   [MAJOR_SPARE] * lay["n_ms"] + [MINOR_SPARE] * lay["n_mi"])
            for k, r in enumerate(self.alive()):
                self.role[r] = seq[k]
            self.pending_advance = False
            self.begin_iteration()
        return self.decision()
