"""CPU oracle for the ZO2 zeroth-order fine-tuning step (test infrastructure only).

Plain, slow, obviously-correct numpy / torch-CPU float64 code written from the
paper (Alg. 1, Alg. 2, Eq. 1-3, Sec. 5.4, Sec. 5.5).  It shares no code with the
HIP library and must never be imported by the product path: only tests, the
smoke check and the bench's cpu_baseline leg may use it.
"""
