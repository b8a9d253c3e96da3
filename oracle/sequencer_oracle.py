"""Plain Python model of the paper's speculative pipelined encryption: test infrastructure.

It follows the paper's description step by step, in its notation, with no cleverness:
  * predictor  f([B_0..B_n], {C_i..C_j}, IV_cur) -> (C_next, IV_next)          (section 5.1)
    patterns: repetitive (weight offloading), FIFO (layer-wise KV swap), LIFO (request-wise);
    predicted IVs carry a leeway for the small transfers that also consume IVs
  * validator  a request matches a pre-encrypted ciphertext when address and length agree and
    the plaintext was not written since                                             (section 5.2)
  * error handler  IV too small -> discard and encrypt now; IV too large -> hold the request
    until the synchronisation and pad NOPs (1-byte transfers that only advance the IV);
    requests inside a batch may be committed in another order than they arrived    (section 5.3)
  * small transfers (below the swap-size threshold) are never pipelined            (section 5.1,
    "Targeting major memory swapping")

The model only decides WHAT happens to which IV; encrypting is somebody else's job.  It emits a
log of actions: ("pre", chunk, iv) encrypt chunk ahead of demand with iv; ("send", chunk, iv)
deliver the pre-encrypted ciphertext; ("now", chunk, iv) encrypt on the critical path and
deliver; ("nop", iv) a 1-byte transfer; ("drop", chunk, iv) discard a pre-encrypted ciphertext.
Only tests may import this module; the C++ sequencer shares nothing with it.
"""

SWAP_THRESHOLD = 128 * 1024     # swaps are usually > 128 KB, other transfers < 8 KB (section 4.2)


class SequencerOracle:
    def __init__(self, iv_start=0, depth=4, leeway=0, threshold=SWAP_THRESHOLD,
                 history_limit=512):
        self.iv_cur = iv_start
        self.depth = depth          # how many future swaps are pre-encrypted
        self.leeway = leeway        # extra IVs left for small transfers between two swaps
        self.threshold = threshold
        self.history_limit = history_limit   # how many past swap-ins the predictor looks at
        self.history = []           # [B_0 .. B_n]: lists of chunks swapped in, batch by batch
        self.batch = []             # the batch being assembled
        self.out = []               # swapped-out chunks not yet swapped in, oldest first
        self.spec = {}              # chunk -> iv of its pre-encrypted ciphertext
        self.pending = []           # requests held until the synchronisation: (chunk, iv)
        self.mode = "fifo"          # which of FIFO / LIFO explained the latest swap-in
        self.log = []

    # ------------------------------------------------------------------ events
    def swap_out(self, chunk):
        """a chunk left the GPU and may come back later"""
        if chunk[1] < self.threshold:
            return                  # small transfers are never pipelined
        if chunk in self.out:
            self.out.remove(chunk)
        self.out.append(chunk)
        self._speculate()

    def notify_write(self, chunk):
        """bytes [address, address + length) changed: every pre-encrypted ciphertext whose
        plaintext range overlaps them is stale (the paper detects this by a page fault)"""
        addr, length = chunk
        served = False
        for c, v in sorted(self.spec.items(), key=lambda e: e[1]):
            if c[0] < addr + length and addr < c[0] + c[1]:
                del self.spec[c]
                self.log.append(("drop", c, v))
                if any(pc == c for pc, _ in self.pending):
                    # a held request loses its ciphertext: it is served on the spot instead
                    self.pending = [(pc, iv) for (pc, iv) in self.pending if pc != c]
                    self.log.append(("now", c, self.iv_cur))
                    self.iv_cur += 1
                    served = True
        if served:
            self._release_pending()
            self._drop_stale()
        self._speculate()

    def request(self, chunk):
        """the application asks for `chunk` = (address, length) to be transferred"""
        addr, length = chunk
        if length < self.threshold:
            # small transfer: encrypted on the spot with the current IV, which may bring the IV
            # to that of a held request
            self.log.append(("now", chunk, self.iv_cur))
            self.iv_cur += 1
            self._release_pending()
            self._drop_stale()
            return
        self._note_swap_in(chunk)
        iv = self.spec.get(chunk)
        if any(chunk == pc for pc, _ in self.pending):
            iv = None               # asked for twice in one batch: the second copy is made now
        if iv is None or iv < self.iv_cur:
            # wrong prediction (or a ciphertext whose IV has passed): relinquish the pipeline,
            # serve the request on the critical path, restart from the ground truth
            for c, v in sorted(self.spec.items(), key=lambda e: e[1]):
                if not any(c == pc for pc, _ in self.pending):
                    self.log.append(("drop", c, v))
            self.spec = {c: v for c, v in self.spec.items()
                         if any(c == pc for pc, _ in self.pending)}
            self.log.append(("now", chunk, self.iv_cur))
            self.iv_cur += 1
            self._release_pending()
            self._drop_stale()
        elif iv == self.iv_cur:
            del self.spec[chunk]
            self.log.append(("send", chunk, iv))
            self.iv_cur += 1
            self._release_pending()
        else:
            # pre-encrypted for a later IV: hold it, another request of the batch may fill the gap
            self.pending.append((chunk, iv))
        self._speculate()

    def sync(self):
        """end of a batch: held requests whose IV still lies ahead are committed in IV order,
        NOPs fill the gaps (inside a batch the order is free: swap re-ordering); those whose IV
        the transfers of the batch have passed are encrypted afresh after them"""
        ahead = sorted((e for e in self.pending if e[1] >= self.iv_cur), key=lambda e: e[1])
        passed = sorted((e for e in self.pending if e[1] < self.iv_cur), key=lambda e: e[1])
        for chunk, iv in ahead:
            while self.iv_cur < iv:
                self.log.append(("nop", self.iv_cur))
                self.iv_cur += 1
            del self.spec[chunk]
            self.log.append(("send", chunk, iv))
            self.iv_cur += 1
        for chunk, iv in passed:
            self.spec.pop(chunk, None)
            self.log.append(("drop", chunk, iv))
            self.log.append(("now", chunk, self.iv_cur))
            self.iv_cur += 1
        self.pending = []
        self._drop_stale()
        if self.batch:
            self.history.append(self.batch)
            self.batch = []
        self._speculate()

    # ------------------------------------------------------------------ internals
    def _release_pending(self):
        """a commit may have advanced the IV to that of a held request"""
        moved = True
        while moved:
            moved = False
            for chunk, iv in list(self.pending):
                if iv == self.iv_cur:
                    self.pending.remove((chunk, iv))
                    del self.spec[chunk]
                    self.log.append(("send", chunk, iv))
                    self.iv_cur += 1
                    moved = True

    def _drop_stale(self):
        """pre-encrypted ciphertexts whose IV lies in the past can never be used"""
        held = {c for c, _ in self.pending}
        for c, v in sorted(self.spec.items(), key=lambda e: e[1]):
            if v < self.iv_cur and c not in held:
                del self.spec[c]
                self.log.append(("drop", c, v))

    def _note_swap_in(self, chunk):
        self.batch.append(chunk)
        if chunk in self.out:
            # which end of the swapped-out set did the application take?
            if len(self.out) > 1:
                if chunk == self.out[0]:
                    self.mode = "fifo"
                elif chunk == self.out[-1]:
                    self.mode = "lifo"
            self.out.remove(chunk)

    def _flat_history(self):
        flat = [c for b in self.history for c in b] + self.batch
        return flat[-self.history_limit:]

    def _predict(self, flat, out, taken):
        """f: the next chunk to be swapped in, or None"""
        # repetitive pattern: the most recent chunk was seen before -> what followed it then
        if flat:
            last = flat[-1]
            for k in range(len(flat) - 2, -1, -1):
                if flat[k] == last:
                    nxt = flat[k + 1]
                    if nxt not in taken:
                        return nxt
                    break
        candidates = [c for c in out if c not in taken]
        if not candidates:
            return None
        return candidates[0] if self.mode == "fifo" else candidates[-1]

    def _speculate(self):
        """keep `depth` predicted swaps pre-encrypted, each with the IV it is expected to meet"""
        # what is already pre-encrypted is the predicted near future: predictions continue from it
        flat = self._flat_history() + [c for c, _ in sorted(self.spec.items(), key=lambda e: e[1])]
        out = [c for c in self.out if c not in self.spec]
        taken = set(self.spec)
        # IVs already promised to pre-encrypted chunks are not reused
        next_iv = max([self.iv_cur] + [v + 1 for v in self.spec.values()])
        while len(self.spec) < self.depth:
            chunk = self._predict(flat, out, taken)
            if chunk is None:
                break
            iv = next_iv + self.leeway
            self.spec[chunk] = iv
            self.log.append(("pre", chunk, iv))
            taken.add(chunk)
            flat = flat + [chunk]
            if chunk in out:
                out.remove(chunk)
            next_iv = iv + 1
