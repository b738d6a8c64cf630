"""CPU oracle for memory-efficient LSTM back-propagation through time.

TEST INFRASTRUCTURE ONLY.  Plain, slow, obviously-correct implementations written from the
paper: the checkpoint-policy dynamic programs, a symbolic executor that counts operations and
checks memory occupancy, and store-everything LSTM BPTT in float64.  Nothing here is used by
the product path, and nothing here imports the HIP library.
"""
