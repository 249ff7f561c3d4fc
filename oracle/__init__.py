"""CPU oracle of the Encode stage (paper section 3.1, Eq. 1).  Test infrastructure only:
imported by tests/, the smoke check and the bench's CPU-baseline leg, never by the
product path."""
