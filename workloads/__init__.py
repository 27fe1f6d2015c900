"""Seeded synthetic inputs shared by the oracle's tests and the GPU path's tests.
Holds random-number recipes only: none of the method's arithmetic lives here."""
